"""MI355X (gfx950) hot path of Independent Subnet Training behind a C ABI.

`ISTContext.partition`, `.subnet_steps` and `.merge` marshal arguments for
ist_partition, ist_subnet_steps and ist_merge of include/ist.h.
"""
from .binding import (EXPORTS, IST_BF16, IST_CSR, IST_DENSE, IST_F32, ISTContext, ISTError,
                      LIB_PATH, load_library, version)


def ist_partition(ctx: ISTContext, Ws, bs, perms, stream=None):
    return ctx.partition(Ws, bs, perms, stream=stream)


def ist_subnet_steps(ctx: ISTContext, y, lr, k, B, X=None, csr=None, **kw):
    return ctx.subnet_steps(y, lr, k, B, X=X, csr=csr, **kw)


def ist_merge(ctx: ISTContext, Ws, bs, stream=None):
    return ctx.merge(Ws, bs, stream=stream)


__all__ = ["ISTContext", "ISTError", "ist_partition", "ist_subnet_steps", "ist_merge",
           "load_library", "version", "EXPORTS", "LIB_PATH"]
