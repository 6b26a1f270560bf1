"""Shared test plumbing: golden loading and trace assembly (no policy arithmetic)."""
import json
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def load_golden(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return json.load(f)


def events_to_arrays(events):
    """[[time, kind, session, dur], ...] -> (ev_time, ev_dur, ev_sk) int32 arrays."""
    ev = np.asarray(events, dtype=np.int64).reshape(-1, 4)
    return (ev[:, 0].astype(np.int32), ev[:, 3].astype(np.int32),
            (ev[:, 2] | (ev[:, 1] << 24)).astype(np.int32))


def code_of(time, outcome, session, slot, host):
    return host | (slot << 10) | (outcome << 12) | (session << 16) | (time << 32)


def digest_of(codes):
    d = 0xCBF29CE484222325
    for c in codes:
        d = (d * 0x100000001B3 + int(c)) & 0xFFFFFFFFFFFFFFFF
    return d
