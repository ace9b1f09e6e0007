"""MI355X-native batched articulated rigid-body simulator (HIP, gfx950).

Thin Python binding over the C ABI declared in include/sim.h: argument
marshalling only, every step of the path runs in the HIP kernels of
libsim355.so.  PyTorch supplies device memory and the stream, nothing else.
"""
from .binding import (Sim, SimError, lib, load_library, CONTACT_DTYPE, PAIR_CONTACT_DTYPE, sim_get_pair_contacts,
                      sim_workspace_bytes, sim_create, sim_create_static, sim_destroy, sim_reset, sim_step, sim_step_obs,
                      sim_get_obs, sim_set_task, sim_get_task_state, sim_get_kept_impulses, sim_set_task_state, sim_set_targets, sim_get_state, sim_set_state,
                      sim_set_step_count, sim_record_contacts, sim_get_contacts,
                      sim_generate_contacts, sim_regroup, sim_set_groups, sim_get_groups, sim_count_near_pairs, sim_check, sim_launch_info, sim_set_envs_per_block, sim_last_error,
                      make_desc, sim_default_params, sim_builtin_robot, SIM_ROBOT_ANT, SIM_ROBOT_HUMANOID)

__all__ = [
    "Sim", "SimError", "lib", "load_library", "CONTACT_DTYPE", "PAIR_CONTACT_DTYPE", "sim_get_pair_contacts", "make_desc",
    "sim_workspace_bytes", "sim_create", "sim_create_static", "sim_destroy", "sim_reset", "sim_step", "sim_step_obs", "sim_get_obs", "sim_set_task", "sim_get_task_state", "sim_get_kept_impulses", "sim_set_task_state",
    "sim_set_targets", "sim_get_state", "sim_set_state", "sim_set_step_count",
    "sim_record_contacts", "sim_get_contacts", "sim_generate_contacts", "sim_regroup", "sim_set_groups", "sim_get_groups", "sim_count_near_pairs", "sim_check",
    "sim_launch_info", "sim_set_envs_per_block", "sim_last_error",
    "sim_default_params", "sim_builtin_robot", "SIM_ROBOT_ANT", "SIM_ROBOT_HUMANOID",
]
