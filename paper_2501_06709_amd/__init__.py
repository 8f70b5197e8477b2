"""MI355X-native paged-KV-cache migration (data path of Mell's adaptive request
migration, arXiv 2501.06709): a thin binding over the C-ABI library libkvm.so.

The names mirror ``include/kvm.h``.  Nothing here computes: pack, unpack, fused
migrate and paged decode all run in the library's HIP kernels.
"""
from .binding import (KVM_BEST_FIT, KVM_BF16, KVM_CLASS_DEFER, KVM_CLASS_KV, KVM_CLASS_TOKENS,
                      KVM_FIRST_FIT, KVM_EHIP, KVM_EINVAL, KVM_ENOMEM, KVM_F16, KVM_OK, Batch, FreeList,
                      KvmError, Pool, kvm_block_bytes, kvm_bytes_per_token,
                      kvm_decode_workspace_bytes, kvm_divide_moves, kvm_layout, kvm_layout_canonical, kvm_migrate,
                      kvm_pack, kvm_paged_decode, kvm_paged_decode_rows, kvm_paged_decode_static, kvm_pool_span_bytes,
                      KVM_STATIC_SCRATCH_BYTES, kvm_set_option,
                      kvm_staging_bytes, kvm_unpack, lib)

__all__ = [n for n in dir() if n.startswith(("kvm_", "KVM_")) or n in
           ("Batch", "FreeList", "KvmError", "Pool", "lib")]
