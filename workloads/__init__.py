"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This package holds data only: kernel templates, launch records, timelines,
page-content generators and the round-robin driver that feeds a memory
scheduler implementation.  None of the method's arithmetic (template
expansion, next-use, victim selection, migration) lives here.
"""
from .trace import (RULE_FIXED, RULE_LINEAR, RULE_STRIDED, RULE_LIST, MAX_ARGS,
                    Rule, Trace, TaskCommands)
from .generators import make_trace, CONFIG_NAMES
from .content import mix64, page_words, stamp_of
from .harness import run_schedule, run_priority_schedule, SwitchRecord

__all__ = [
    "RULE_FIXED", "RULE_LINEAR", "RULE_STRIDED", "RULE_LIST", "MAX_ARGS",
    "Rule", "Trace", "TaskCommands", "make_trace", "CONFIG_NAMES",
    "mix64", "page_words", "stamp_of", "run_schedule", "run_priority_schedule", "SwitchRecord",
]
