"""CPU oracle for the bounded self-speculative decode step.

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's cpu_baseline leg.  The HIP library never imports or calls it, and it
never imports the HIP library.
"""
from .oracle import (Oracle, OracleSession, OrcParams, load_lib, matvec, rmsnorm, swiglu, act,
                     rope_angles, rope_apply, attention_head, sample_dist, sample_token, temperature_schedule,
                     expected_accept, round_time, speedup, EXITED, WIDTH_BOUND, DEPTH_BOUND,
                     PH_DRAFT, PH_ALIGN, PH_VERIFY, num_threads)

__all__ = ["Oracle", "OracleSession", "OrcParams", "load_lib", "matvec", "rmsnorm", "swiglu", "act",
           "rope_angles", "rope_apply", "attention_head", "sample_dist", "sample_token", "temperature_schedule",
           "expected_accept", "round_time", "speedup", "EXITED", "WIDTH_BOUND",
           "DEPTH_BOUND", "PH_DRAFT", "PH_ALIGN", "PH_VERIFY", "num_threads"]
