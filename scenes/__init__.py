"""Seeded synthetic inputs: robot tables, terrains, env placement, actions, poses.

This module only *describes* workloads (numbers that are handed to a simulator
as input).  It holds none of the simulation step's arithmetic and imports
neither the HIP binding nor the CPU oracle; both are fed from here.

The robots are self-designed stick figures whose sizes sit inside the ranges of
the paper's Ant and Humanoid tasks (Section 4.1: 4 legs / 8 actuated joints, and
28-DoF humanoid with 21 actuated joints); the terrain stands in for the uneven
ground with rectangular obstacles of the complex-terrain task.
"""
from .robots import (Robot, make_ant, make_humanoid, make_chain, make_single, make_star, make_raft, make_loose,
                     capsule_mass_inertia, collision_pairs, LOCK, HINGE)
from .terrain import (Terrain, make_plane, make_heightfield, make_flat_heightfield,
                      make_tilted_heightfield, terrain_height_max_near, PLANE, HEIGHTFIELD)
from .workloads import (Scene, SimParams, TaskParams, make_scene, config_scene, crowd_origins, CONFIGS,
                        actions_for_step, targets_for_step, fallen_states, rest_state,
                        posed_state, env_grid_origins)

__all__ = [
    "Robot", "make_ant", "make_humanoid", "make_chain", "make_single", "make_star", "make_raft", "make_loose",
    "capsule_mass_inertia", "collision_pairs",
    "LOCK", "HINGE", "Terrain", "make_plane", "make_heightfield", "make_flat_heightfield",
    "make_tilted_heightfield", "terrain_height_max_near", "PLANE", "HEIGHTFIELD",
    "Scene", "SimParams", "TaskParams", "make_scene", "config_scene", "crowd_origins", "CONFIGS",
    "actions_for_step", "targets_for_step", "fallen_states", "rest_state", "posed_state",
    "env_grid_origins",
]
