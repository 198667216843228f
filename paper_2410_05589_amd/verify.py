"""ctypes binding of the tree-construction and acceptance-walk entry points (include/ps_verify.h):
same names as the C ABI, argument marshalling only; the work runs in the HIP library."""
import ctypes

import numpy as np

from . import binding as B

PS_TREE_MAX_NODES = 64
EXPORTED_SYMBOLS = ("ps_tree_tokens", "ps_verify_walk", "ps_verify_workspace_bytes", "ps_verify_walk_static")


class ps_tree_shape(ctypes.Structure):
    _fields_ = [("n_nodes", ctypes.c_int32), ("parent", ctypes.POINTER(ctypes.c_int32)),
                ("rank", ctypes.POINTER(ctypes.c_int32))]


class ps_verify_args(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("rows", ctypes.c_int32), ("vocab", ctypes.c_int32),
                ("tokens", ctypes.c_void_p), ("q", ctypes.c_void_p), ("p", ctypes.c_void_p), ("r", ctypes.c_void_p),
                ("n_accepted", ctypes.c_void_p), ("path", ctypes.c_void_p),
                ("out_tokens", ctypes.c_void_p), ("top_ids", ctypes.c_void_p), ("topk", ctypes.c_int32),
                ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t)]


_ready = False


def _lib():
    global _ready
    lib = B.load_library()
    if not _ready:
        lib.ps_tree_tokens.restype = ctypes.c_int
        lib.ps_tree_tokens.argtypes = [ctypes.POINTER(ps_tree_shape), ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                       ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.ps_verify_walk.restype = ctypes.c_int
        lib.ps_verify_walk.argtypes = [ctypes.POINTER(ps_tree_shape), ctypes.POINTER(ps_verify_args), ctypes.c_void_p]
        lib.ps_verify_walk_static.restype = ctypes.c_int
        lib.ps_verify_walk_static.argtypes = lib.ps_verify_walk.argtypes
        lib.ps_verify_workspace_bytes.restype = ctypes.c_size_t
        lib.ps_verify_workspace_bytes.argtypes = [ctypes.c_int32, ctypes.c_int32]
        _ready = True
    return lib


def make_tree(parent, rank=None):
    """ps_tree_shape over host arrays (kept alive by the returned object)."""
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    t = ps_tree_shape()
    t.n_nodes = len(parent)
    t._parent = parent
    t.parent = parent.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    if rank is not None:
        rank = np.ascontiguousarray(rank, dtype=np.int32)
        assert len(rank) == len(parent)
        t._rank = rank
        t.rank = rank.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    return t


def ps_tree_tokens(tree, batch, rows, topk, top_ids_ptr, tokens_ptr, stream_ptr):
    return _lib().ps_tree_tokens(ctypes.byref(tree) if tree is not None else None, batch, rows, topk,
                                 top_ids_ptr, tokens_ptr, stream_ptr)


def ps_verify_walk(tree, args, stream_ptr):
    return _lib().ps_verify_walk(ctypes.byref(tree) if tree is not None else None,
                                 ctypes.byref(args) if args is not None else None, stream_ptr)


def ps_verify_walk_static(tree, args, stream_ptr):
    return _lib().ps_verify_walk_static(ctypes.byref(tree) if tree is not None else None,
                                        ctypes.byref(args) if args is not None else None, stream_ptr)


def ps_verify_workspace_bytes(batch, vocab):
    return int(_lib().ps_verify_workspace_bytes(batch, vocab))
