# placeholder until the C-ABI library exists
class PowerAttnError(RuntimeError):
    pass
def library_path(): raise PowerAttnError("not built")
def load_library(): raise PowerAttnError("not built")
def power_attn_fwd(*a, **k): raise PowerAttnError("not built")
def power_attn_bwd(*a, **k): raise PowerAttnError("not built")
def power_attn_workspace_bytes(*a, **k): raise PowerAttnError("not built")
