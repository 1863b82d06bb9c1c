"""MI355X-native forward pass of CNN blocks in the original and slim forms of DeepRebirth.

``binding``  - ctypes access to the C ABI of libdeeprebirth.so (the only compute path)
``graph``    - layer lists -> library descriptors / device parameters
``slim``     - streamline and branch slimming as transforms on layer lists
``build``    - compiles the library for gfx950
"""
