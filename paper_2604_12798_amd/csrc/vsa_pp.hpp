// Host-side entry points of vsa_pp.hip (internal to libvfa.so; not part of the C ABI in vfa.h).  The kernel parameter
// block is a type of an anonymous namespace, so it crosses the translation-unit boundary as bytes.
#pragma once

#pragma GCC visibility push(hidden)
// hipFuncSetAttribute(max dynamic LDS) for attn_vsa_pp_kernel on the current device; 0 on success
int vfa_detail_vsa_pp_raise_lds(void);
// launches attn_vsa_pp_kernel with n_wg workgroups of 512 threads on `stream`; `params` points to a Params object of
// `params_bytes` bytes; 0 on success
int vfa_detail_vsa_pp_launch(const void* params, unsigned long params_bytes, unsigned n_wg, void* stream);
#pragma GCC visibility pop
