"""MI355X-native AdaDim layer search (ctypes binding is loaded lazily)."""
