"""Runs the host-side test files against AddressSanitizer + UBSan builds of the library's
planner and of the C checker.  Started by test_sanitized_host.py in a process of its own
with the sanitizer runtime preloaded; not collected by pytest (no test_ prefix).

usage: sanitized_runner.py <planner .so> <checker .so>"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(HERE))
sys.path.insert(0, HERE)

# the planner's host entry points: everything planner.cpp defines, nothing that launches
HOST_ONLY = ("craft_status_str", "craft_plan", "craft_plan_destroy", "craft_plan_summary",
             "craft_plan_layer_info", "craft_plan_layer_tables", "craft_plan_greedy_order",
             "craft_plan_benefit", "craft_plan_rank_rows", "craft_plan_diff", "craft_plan_tables_bytes")


def main():
    planner_so, checker_so = sys.argv[1], sys.argv[2]
    import pytest
    import oracle
    from paper_2603_28768_amd import binding
    oracle._LIB = checker_so
    oracle.build = lambda force=False: checker_so                  # already built, with the sanitizers
    binding.LIB_PATH = planner_so
    binding.EXPORTS = {k: v for k, v in binding.EXPORTS.items() if k in HOST_ONLY}
    # tests that need device entry points (workspace and tile queries live beside the launches)
    skip = "not tile_heights and not workspace_query and not static_scratch and not argument_checks"
    files = [os.path.join(HERE, f) for f in ("test_plan_host.py", "test_oracle_forward.py", "test_oracle_e4m3.py",
                                             "test_oracle_router_logits.py")]
    return pytest.main(["-x", "-q", "-p", "no:cacheprovider", "-k", skip, *files])


if __name__ == "__main__":
    sys.exit(main())
