"""Seeded synthetic inputs for the LOMO hot path (shapes of LLaMA 7B/13B/65B layers).

This module only *makes inputs*: fp16 tensors, token ids and the five workload
descriptions.  It contains none of the method's arithmetic (no gradients, norms,
updates) and is the only code that both the CPU oracle's tests and the HIP path's
tests share.  Every generator is counter based, so any row/column subset of a
tensor can be produced on the CPU without generating the whole tensor, and the
device twin (torch integer ops, used as plumbing) yields the same bits.
"""
from .generators import (tensor_key, normal_f16_np, normal_f16_torch, normal_mult,
                         zipf_ids, splitmix64_np)
from .configs import (TensorSpec, Workload, workload, llama_tensor_list, WORKLOAD_NAMES,
                      count_params, StreamedStack)

__all__ = ["tensor_key", "normal_f16_np", "normal_f16_torch", "normal_mult", "zipf_ids",
           "splitmix64_np", "TensorSpec", "Workload", "workload", "llama_tensor_list",
           "WORKLOAD_NAMES", "count_params", "StreamedStack"]
