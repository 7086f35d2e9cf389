"""The host-only rows (sampler partition, online re-planning, two-level
weights, share planning, bucket layout) checked against the CPU checker with
the library as it is loaded on the GPU machine: the same property checks that
run without a GPU, re-run under the `gpu` marker so that a GPU test run covers
every entry point of the library it loads."""
import sys

import pytest

import test_host_api as host_api

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def announce(request):
    print("\n[gpu-case] %s" % request.node.nodeid, file=sys.stderr, flush=True)
    yield


def test_sampler_partition_on_the_gpu_machine():
    host_api.test_sampler_bit_exact_vs_checker()
    host_api.test_sampler_paper_setting_and_errors()


def test_online_replanning_on_the_gpu_machine():
    host_api.test_replan_bit_exact_vs_checker()
    host_api.test_replan_errors_leave_state_untouched()


def test_two_level_weights_on_the_gpu_machine():
    host_api.test_group_weights_bit_exact_vs_checker()
    host_api.test_group_weights_errors()


def test_shares_and_layout_on_the_gpu_machine():
    host_api.test_shares_bit_exact_vs_checker()
    host_api.test_shares_workloads_and_golden()
    host_api.test_layout_and_tiles_vs_checker()
    host_api.test_layout_workloads_vs_checker()
