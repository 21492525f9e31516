THI_OK=0
class ThiError(RuntimeError): pass
class Workspace: pass
def library_path(): pass
def load_library(): pass
def thi_linear(*a): pass
def thi_rmsnorm_qkv(*a): pass
def thi_swiglu_mlp(*a): pass
def thi_status_string(*a): pass
def thi_version(): pass
def thi_workspace_bytes(*a): pass
def thi_workspace_init(*a): pass
