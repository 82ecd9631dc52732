"""Host logic of the library run on the GPU machine as well (the same checks the CPU tier runs): the planner's
C-ABI entry points against the Python reference, and the launch-grouping query."""
import pytest

pytestmark = pytest.mark.gpu


def test_planner_parity_on_the_gpu_box():
    import test_planner_parity as t
    t.test_table8_workload()
    t.test_random_problems_agree()
    t.test_bad_inputs_are_rejected()
    t.test_strategy_table_with_the_r3_curve_measured_on_mi355x()


def test_pipeline_query_on_the_gpu_box():
    import test_abi_host as t
    t.test_pipeline_query_reports_the_launch_grouping()
