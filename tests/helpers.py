"""Re-export of the oracle-side plumbing for the tests."""
from oracle.packs import (compact_packs, compact_weights, dense_packs, err_metric, key_valid_of,  # noqa: F401
                          oracle_masks)


def make_wl(spec, **kw):
    """A synthetic workload with the ORACLE's key mask attached as `key_valid` (the library derives its own on the
    device from the same presence masks; test_key_valid_matches_oracle compares the two)."""
    from paper_2604_08971_amd import workloads as W
    wl = W.make_workload(spec, **kw)
    wl.key_valid = key_valid_of(wl)
    return wl
