"""MI355X-native SkipKV compression step (score -> select -> compact, steering add).

Importing the package loads nothing native; `paper_2512_07993_amd.binding` loads
libskipkv.so on first use and raises if it has not been built.
"""
__version__ = "0.1.0"
